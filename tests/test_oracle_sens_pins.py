"""Pins for the oracle's per-scenario stage times and link sensitivities: an explicit
dependency graph solved by networkx, the closed forms of the absorbed and the cascading
regime (Theorem 1, Eq. (1)), and structural properties.  No GPU needed."""
import networkx as nx
import numpy as np

from test_oracle_pins import build_dag, rand_instance

INT32_MAX = 2 ** 31 - 1


def _dag_makespan(S, M, t_f, t_b, w, cf, cb):
    G, _ = build_dag(S, M, t_f, t_b, w, cf, cb)
    return nx.dag_longest_path_length(G, weight="weight")


def test_sensitivity_equals_dag_longest_path_differences(oracle):
    rng = np.random.default_rng(4242)
    for trial in range(25):
        S, M = int(rng.integers(2, 6)), int(rng.integers(2, 9))
        t_f, t_b, w, cf, cb = rand_instance(rng, S, M, valid=True, c_hi=60)
        delta = int(rng.integers(1, 40))
        r = oracle.sensitivity(S, M, t_f, t_b, np.full(S, M + 1), w[:, None], cf[:, None], cb[:, None], delta)
        base = _dag_makespan(S, M, t_f, t_b, w, cf, cb)
        assert r["makespan"][0, 0] == base
        for l in range(S - 1):
            up = cf.copy()
            up[l] += delta
            assert r["sens"][0, l, 0] == _dag_makespan(S, M, t_f, t_b, w, up, cb) - base, (trial, l)


def test_per_scenario_stage_times_equal_dag_longest_path(oracle):
    rng = np.random.default_rng(777)
    S, M, K, C = 4, 6, 5, 3
    tfs = rng.integers(1, 60, (S, K))
    tbs = rng.integers(1, 90, (S, K))
    cf = rng.integers(0, 100, (S - 1, K))
    cb = rng.integers(0, 100, (S - 1, K))
    w = np.sort(rng.integers(0, M, (S, C)), axis=0)[::-1].copy()
    r = oracle.eval_scenario_times(S, M, tfs, tbs, np.full(S, M + 1), w, cf, cb)
    assert r["makespan"].shape == (K, C) and r["bubble"].shape == (S, K, C)
    for k in range(K):
        for c in range(C):
            mk = _dag_makespan(S, M, tfs[:, k], tbs[:, k], w[:, c], cf[:, k], cb[:, k])
            assert r["makespan"][k, c] == mk
            for s in range(S):
                assert r["bubble"][s, k, c] == mk - M * (tfs[s, k] + tbs[s, k])


def test_absorbed_regime_every_link_costs_exactly_delta(oracle):
    """Uniform stage times with Eq. (1) true on every link, before and after the
    perturbation: makespan = (M+S-1)(t_f+t_b) + all link delays, so each link's finite
    difference is exactly delta (the one-off lead-in) -- never more."""
    rng = np.random.default_rng(31)
    hits = 0
    for _ in range(200):
        S, M = int(rng.integers(2, 7)), int(rng.integers(10, 40))
        tf, tb = int(rng.integers(2, 40)), int(rng.integers(2, 40))
        tau = tf + tb
        d = rng.integers(2, 4, S - 1)
        w = np.concatenate([np.cumsum(d[::-1])[::-1], [0]])
        if w[0] > M - 1:
            continue
        delta = int(rng.integers(1, tau + 1))
        cf = np.array([rng.integers(0, (x - 1) * tau - delta + 1) for x in d])
        cb = np.array([rng.integers(0, (x - 1) * tau - delta - cf[i] + 1) for i, x in enumerate(d)])
        r = oracle.sensitivity(S, M, np.full(S, tf), np.full(S, tb), np.full(S, M + 1),
                               w[:, None], cf[:, None], cb[:, None], delta)
        assert np.all(r["sens"] == delta)
        hits += 1
    assert hits > 50


def test_cascading_regime_pays_delta_once_per_group(oracle):
    """Theorem 1, uniform times t, slack Delta on one link whose delay c > (Delta-1) t each
    way: every Delta+1 further micro-batches cost 4t + c_fwd + c_bwd, so raising c_fwd by
    delta costs delta once per group -- the finite difference grows by n delta over n
    groups, while an absorbing link's stays put."""
    S, t, link, Delta = 4, 10, 1, 2
    t_f = t_b = np.full(S, t)
    w = np.zeros(S, dtype=np.int64)
    for s in range(S - 2, -1, -1):
        w[s] = w[s + 1] + (Delta if s == link else 1)
    cf = np.zeros((S - 1, 1), dtype=np.int64)
    cf[link] = 3 * t
    cb = cf.copy()
    delta, n, M0 = 7, 9, 40
    a = oracle.sensitivity(S, M0, t_f, t_b, np.full(S, 10 ** 6), w[:, None], cf, cb, delta)["sens"][0, :, 0]
    b = oracle.sensitivity(S, M0 + n * (Delta + 1), t_f, t_b, np.full(S, 10 ** 6), w[:, None], cf, cb, delta)["sens"][0, :, 0]
    assert b[link] - a[link] == n * delta
    assert a[link] > delta
    for l in range(S - 1):
        if l != link:
            assert a[l] == b[l]


def test_hidden_link_has_zero_sensitivity(oracle):
    """Stage 0 far slower than the rest and enough warm-up forwards: stage 0 never waits, the
    makespan is M (t_f[0] + t_b[0]) and no link delay is on the critical path."""
    S, M = 4, 24
    t_f = np.array([100, 5, 5, 5])
    t_b = np.array([200, 5, 5, 5])
    w = np.array([6, 2, 1, 0])
    cf = np.full((S - 1, 1), 20)
    cb = np.full((S - 1, 1), 20)
    r = oracle.sensitivity(S, M, t_f, t_b, np.full(S, M + 1), w[:, None], cf, cb, 15)
    assert r["makespan"][0, 0] == M * 300
    assert np.all(r["sens"] == 0)


def test_makespan_depends_on_a_link_only_through_its_round_trip(oracle):
    """Moving delay between the two directions of a link shifts the downstream stages'
    timelines but not the makespan, so forward and backward sensitivities coincide (the
    paper's Eq. (1) sees a link through 2 c_i only)."""
    rng = np.random.default_rng(99)
    for _ in range(20):
        S, M = int(rng.integers(2, 7)), int(rng.integers(2, 14))
        t_f, t_b, w, cf, cb = rand_instance(rng, S, M, valid=True, c_hi=80)
        delta = int(rng.integers(1, 50))
        args = (S, M, t_f, t_b, np.full(S, M + 1), w[:, None], cf[:, None], cb[:, None], delta)
        f = oracle.sensitivity(*args, direction="fwd")
        b = oracle.sensitivity(*args, direction="bwd")
        assert np.array_equal(f["sens"], b["sens"])
        tot = cf + cb
        moved = oracle.sensitivity(S, M, t_f, t_b, np.full(S, M + 1), w[:, None],
                                   tot[:, None], np.zeros((S - 1, 1), dtype=np.int64), delta)
        assert np.array_equal(moved["makespan"], f["makespan"])


def test_deadlocked_candidate_gets_sentinels(oracle):
    S, M = 3, 5
    w = np.array([[2, 0], [1, 2], [0, 1]])          # candidate 1 violates Lemma 1
    r = oracle.sensitivity(S, M, np.full(S, 3), np.full(S, 4), np.full(S, M + 1), w,
                           np.ones((S - 1, 2), dtype=np.int64), np.ones((S - 1, 2), dtype=np.int64), 2)
    assert np.all(r["sens"][1] == INT32_MAX) and np.all(r["makespan"][1] == INT32_MAX)
    assert np.all(r["sens"][0] < INT32_MAX)
