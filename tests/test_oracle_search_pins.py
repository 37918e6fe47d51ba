"""Pins for the oracle's guided search: a descent worked by hand from the closed forms of
Theorem 1 / Eq. (1), local optimality by direct enumeration of the neighbourhood, and bounds
against the exhaustive optimum.  No GPU needed."""
import itertools

import numpy as np
import pytest

from oracle import search as osearch

INT32_MAX = 2 ** 31 - 1


def test_hand_worked_descent_two_stages(oracle):
    """S = 2, t_f = t_b = 10 on both stages, 25 us each way on the link.  Eq. (1) asks for
    20 + 50 <= Delta 20, i.e. Delta >= 4.  Below that every group of Delta + 1 micro-batches
    pays 4t + 2c (Theorem 1), so each +1 on Delta is a strict gain; from Delta = 4 on the makespan
    is (M + S - 1) 20 + 50 and nothing improves.  From w = (1, 0): three moving rounds
    (the first prices the start and its neighbours and goes to Delta 2, then 3, then 4) and a
    fourth that finds nothing."""
    S, M = 2, 60
    t = np.full(S, 10)
    cf = np.full((1, 1), 25)
    for nb in (0, 1):
        r = osearch.search(S, M, t, t, np.full(S, M), np.array([1, 0]), cf, cf, neighbourhood=nb)
        assert list(r["w"][:, 0]) == [4, 0]
        assert r["makespan"][0] == (M + S - 1) * 20 + 50
        assert r["rounds"] == 4


def test_memory_cap_stops_the_descent(oracle):
    """Same pipeline, but stage 0 may hold 3 activations (x_0 = w_0 + 1 <= 3): the descent stops
    at Delta = 2, a point the closed form of the cascading regime prices."""
    S, M = 2, 60
    t = np.full(S, 10)
    cf = np.full((1, 1), 25)
    r = osearch.search(S, M, t, t, np.array([3, 3]), np.array([1, 0]), cf, cf, neighbourhood=0)
    assert list(r["w"][:, 0]) == [2, 0]
    assert r["rounds"] == 2
    tl = oracle.timeline(S, M, t, t, np.array([2, 0]), cf[:, 0], cf[:, 0])
    assert r["makespan"][0] == tl["makespan"]


def test_move_lists():
    assert osearch.moves(3, 0) == [(0, 0, -1), (0, 0, 1), (0, 1, -1), (0, 1, 1), (0, 2, -1), (0, 2, 1)]
    m1 = osearch.moves(3, 1)
    assert len(m1) == 3 * 4 and m1[:4] == [(0, 0, -1), (0, 0, 1), (0, 1, -1), (0, 1, 1)]
    assert set(osearch.moves(4, 0)) <= set(osearch.moves(4, 1))


def _makespan_or_none(oracle, S, M, t_f, t_b, cap, w, cf, cb):
    """Feasible makespan from the timeline routine (a different entry of the simulator than the
    one the search uses), None if Lemma 1 or the cap rules the vector out."""
    if any(w[s] < w[s + 1] for s in range(S - 1)) or any(w[s] + 1 > cap[s] for s in range(S)):
        return None
    return oracle.timeline(S, M, t_f, t_b, w, cf, cb)["makespan"]


@pytest.mark.parametrize("nb", [0, 1])
def test_result_is_a_local_optimum_and_bounded_by_the_exhaustive_one(oracle, nb):
    rng = np.random.default_rng(2024 + nb)
    reached = total = 0
    for trial in range(12):
        S, M, K = int(rng.integers(2, 5)), int(rng.integers(6, 12)), 6
        t_f = rng.integers(5, 30, S)
        t_b = rng.integers(5, 50, S)
        cf = rng.integers(0, 200, (S - 1, K))
        cb = rng.integers(0, 200, (S - 1, K))
        cap = rng.integers(S, M + 1, S)
        cap = np.maximum(cap, np.arange(S, 0, -1))              # plain 1F1B always fits
        start = np.arange(S - 1, -1, -1)
        r = osearch.search(S, M, t_f, t_b, cap, start, cf, cb, neighbourhood=nb)
        assert r["rounds"] >= 1
        for k in range(K):
            w = r["w"][:, k].astype(np.int64)
            here = _makespan_or_none(oracle, S, M, t_f, t_b, cap, w, cf[:, k], cb[:, k])
            assert here is not None and here == r["makespan"][k]
            s0 = _makespan_or_none(oracle, S, M, t_f, t_b, cap, start, cf[:, k], cb[:, k])
            assert here <= s0
            # no move of the neighbourhood improves (own neighbours: a subset of what the pool held)
            for a, b, sign in osearch.moves(S, nb):
                q = w.copy()
                q[a:b + 1] += sign
                q = np.clip(q, 0, M - 1)
                v = _makespan_or_none(oracle, S, M, t_f, t_b, cap, q, cf[:, k], cb[:, k])
                assert v is None or v >= here
            # exhaustive optimum over every vector
            best = min(v for v in (_makespan_or_none(oracle, S, M, t_f, t_b, cap, np.array(q), cf[:, k], cb[:, k])
                                   for q in itertools.product(range(M), repeat=S)) if v is not None)
            assert here >= best
            reached += here == best
            total += 1
    assert reached >= 0.5 * total          # a heuristic, but not a useless one on small pipelines


def test_scenarios_descend_independently(oracle):
    """The result for a scenario is what the search finds on that scenario alone; only the
    number of rounds is shared (the slowest descent's)."""
    rng = np.random.default_rng(77)
    S, M, K = 4, 14, 7
    t_f, t_b = rng.integers(5, 30, S), rng.integers(5, 50, S)
    cf, cb = rng.integers(0, 300, (S - 1, K)), rng.integers(0, 300, (S - 1, K))
    cap = np.full(S, M)
    start = np.arange(S - 1, -1, -1)
    for nb in (0, 1):
        together = osearch.search(S, M, t_f, t_b, cap, start, cf, cb, neighbourhood=nb)
        rounds = []
        for k in range(K):
            alone = osearch.search(S, M, t_f, t_b, cap, start, cf[:, k:k + 1], cb[:, k:k + 1], neighbourhood=nb)
            assert np.array_equal(alone["w"][:, 0], together["w"][:, k])
            assert alone["makespan"][0] == together["makespan"][k]
            rounds.append(alone["rounds"])
        assert together["rounds"] == max(rounds)
        assert together["evaluated"] == together["rounds"] * K * (len(osearch.moves(S, nb)) + 1)


def test_a_scenario_without_delays_stays_where_it_is(oracle):
    S, M = 2, 60
    t = np.full(S, 10)
    z = np.zeros((1, 1), dtype=np.int64)
    alone = osearch.search(S, M, t, t, np.full(S, M), np.array([1, 0]), z, z)
    # round 1 prices the start (its makespan was unknown), round 2 finds nothing better
    assert alone["rounds"] == 2 and list(alone["w"][:, 0]) == [1, 0]
    assert alone["makespan"][0] == (M + S - 1) * 20


def test_infeasible_start_without_feasible_neighbour(oracle):
    S, M = 3, 8
    t = np.full(S, 10)
    cf = np.zeros((S - 1, 2), dtype=np.int64)
    r = osearch.search(S, M, t, t, np.zeros(S, dtype=np.int64), np.array([2, 1, 0]), cf, cf)
    assert np.all(r["makespan"] == INT32_MAX) and r["rounds"] == 1
