"""Pins for the analytic planning oracle (Algorithm 1, Algorithm 2, Eq. (1)): values worked
out by hand from the paper's listings, the optimality the paper claims for Algorithm 1 by
brute force, and the purpose of Algorithm 2 checked on the event-driven simulator."""
import itertools

import numpy as np
import pytest

from oracle import seed


def test_algorithm1_hand_worked_values():
    # S=4, x_max=7: avg = 6 // 3 = 2, r = 0            -> 7 5 3 1
    assert seed.initial_plan(4, 7) == [7, 5, 3, 1]
    # S=4, x_max=8: avg = 7 // 3 = 2, r = 1, link 0 +1 -> 8 5 3 1
    assert seed.initial_plan(4, 8) == [8, 5, 3, 1]
    # S=5, x_max=3: avg = 0, r = 2                     -> 3 2 1 1 1
    assert seed.initial_plan(5, 3) == [3, 2, 1, 1, 1]
    assert seed.initial_plan(1, 6) == [6]
    assert seed.initial_plan(3, 1) == [1, 1, 1]
    # x_max = S is plain 1F1B
    assert seed.to_w(seed.initial_plan(6, 6)) == [5, 4, 3, 2, 1, 0]


@pytest.mark.parametrize("S", [2, 3, 4, 5])
def test_algorithm1_maximises_the_minimum_slack(S):
    """Section 4.2: the initial plan maximises min_i Delta_i under x_0 <= x_max, x_{S-1} >= 1
    and Lemma 1; its slack is as balanced as possible; x_0 = x_max, x_{S-1} = 1."""
    for x_max in range(1, 10):
        x = seed.initial_plan(S, x_max)
        d = [x[i] - x[i + 1] for i in range(S - 1)]
        assert x[0] == x_max and x[-1] == 1
        assert all(v >= 0 for v in d) and max(d) - min(d) <= 1
        best = -1
        for cand in itertools.product(range(1, x_max + 1), repeat=S):
            dd = [cand[i] - cand[i + 1] for i in range(S - 1)]
            if min(dd) >= 0:
                best = max(best, min(dd))
        assert min(d) == best


def test_algorithm2_hand_worked_values():
    # S=3, t_f=10, t_b=20 everywhere, delay 15 both ways on link 0 only, N large:
    # link 1: ceil(30/30) = 1 -> 2, x_1 = 3;  link 0: ceil((30+30)/30) = 2, x_0 = 5
    assert seed.adapted_plan(3, 100, [10] * 3, [20] * 3, [15, 0], [15, 0]) == [5, 3, 1]
    # a slower delay: ceil((30+2*40)/30) = 4
    assert seed.adapted_plan(3, 100, [10] * 3, [20] * 3, [40, 0], [40, 0]) == [7, 3, 1]
    # the clip N - 2S = 3 bites on link 0
    assert seed.adapted_plan(3, 9, [10] * 3, [20] * 3, [400, 0], [400, 0]) == [6, 3, 1]
    # N - 2S = 0: no slack at all; N - 2S < 0 is floored at 0 (Lemma 1)
    assert seed.adapted_plan(4, 8, [10] * 4, [20] * 4, [5] * 3, [5] * 3) == [1, 1, 1, 1]
    assert seed.adapted_plan(4, 6, [10] * 4, [20] * 4, [5] * 3, [5] * 3) == [1, 1, 1, 1]
    # heterogeneous stages: link 1 ceil((8+12+6)/(20+30)) = 1 -> 2; link 0 ceil((50+70+20)/(8+12)) = 7
    assert seed.adapted_plan(3, 64, [50, 8, 20], [70, 12, 30], [10, 3], [10, 3]) == [10, 3, 1]


def test_algorithm2_gives_the_smallest_slack_that_satisfies_eq1():
    rng = np.random.default_rng(3)
    for _ in range(300):
        S = int(rng.integers(2, 9))
        N = 10 ** 6          # neither the clip N - 2S nor the cap x <= N applies
        t_f, t_b = rng.integers(1, 100, S), rng.integers(1, 200, S)
        cf, cb = rng.integers(0, 3000, S - 1), rng.integers(0, 3000, S - 1)
        x = seed.adapted_plan(S, N, t_f, t_b, cf, cb)
        w = seed.to_w(x)
        assert x[-1] == 1 and all(x[i] - x[i + 1] >= 2 for i in range(S - 1))
        assert all(seed.absorbed(S, t_f, t_b, w, cf, cb))
        for i in range(S - 1):
            if x[i] - x[i + 1] > 2:           # one forward less on this link breaks Eq. (1)
                w2 = list(w)
                for j in range(i + 1):
                    w2[j] -= 1
                assert not seed.absorbed(S, t_f, t_b, w2, cf, cb)[i]


def test_algorithm2_schedule_does_not_cascade_on_the_simulator(oracle):
    """What Algorithm 2 is for: with its warm-up counts the delays are absorbed, so every
    further micro-batch costs exactly the slowest stage's t_f + t_b (simulated)."""
    rng = np.random.default_rng(9)
    for _ in range(40):
        S = int(rng.integers(2, 7))
        t_f, t_b = rng.integers(5, 60, S), rng.integers(5, 90, S)
        cf, cb = rng.integers(0, 600, S - 1), rng.integers(0, 600, S - 1)
        w = seed.to_w(seed.adapted_plan(S, 10 ** 6, t_f, t_b, cf, cb))
        M0 = 3 * w[0] + 300                       # well past the transient
        a = oracle.timeline(S, M0, t_f, t_b, w, cf, cb)["makespan"]
        b = oracle.timeline(S, M0 + 25, t_f, t_b, w, cf, cb)["makespan"]
        assert b - a == 25 * int((t_f + t_b).max())
        # ... while plain 1F1B under the same delays does cascade whenever Eq. (1) fails for it
        w1 = list(range(S - 1, -1, -1))
        if not all(seed.absorbed(S, t_f, t_b, w1, cf, cb)):
            a1 = oracle.timeline(S, M0, t_f, t_b, w1, cf, cb)["makespan"]
            b1 = oracle.timeline(S, M0 + 25, t_f, t_b, w1, cf, cb)["makespan"]
            worst = max((int(t_f[i] + t_b[i] + t_f[i + 1] + t_b[i + 1] + cf[i] + cb[i]) + 1) // 2 for i in range(S - 1))
            if worst > int((t_f + t_b).max()):
                assert b1 - a1 > 25 * int((t_f + t_b).max())


def test_eq1_oracle_marks_exactly_the_link_that_cascades(oracle):
    """absorbed() against the simulator: slack 2 everywhere, one slow link; the growth per
    micro-batch stays at the bottleneck stage's period iff absorbed() says so."""
    rng = np.random.default_rng(21)
    S = 5
    for _ in range(60):
        t_f, t_b = rng.integers(5, 30, S), rng.integers(5, 40, S)
        tau = t_f + t_b
        link = int(rng.integers(0, S - 1))
        cf, cb = np.zeros(S - 1, dtype=np.int64), np.zeros(S - 1, dtype=np.int64)
        cf[link], cb[link] = rng.integers(0, 150, 2)
        w = [6 * (S - 1 - s) for s in range(S)]        # ample slack on every other link
        w = [v - (0 if s > link else 4) for s, v in enumerate(w)]      # slack 2 on the slow link
        ok = seed.absorbed(S, t_f, t_b, w, cf, cb)
        assert all(ok[i] for i in range(S - 1) if i != link)
        a = oracle.timeline(S, 900, t_f, t_b, w, cf, cb)["makespan"]       # well past the transient
        b = oracle.timeline(S, 900 + 30, t_f, t_b, w, cf, cb)["makespan"]
        # cycle through the slow link: (tau_i + tau_{i+1} + cf + cb) per Delta + 1 = 3 micro-batches
        cyc = int(tau[link] + tau[link + 1] + cf[link] + cb[link])
        if ok[link]:
            assert cyc <= 3 * int(tau[link + 1])
        if 3 * int(tau.max()) >= cyc:
            assert b - a == 30 * int(tau.max())
        else:
            assert b - a == 10 * cyc and not ok[link]
