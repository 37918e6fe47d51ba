"""Pins for the CPU oracle: everything here checks the event-driven simulator
against something other than itself -- an explicit dependency graph solved by a
library longest-path routine, closed forms, the paper's Lemma 1 / Theorem 1 /
Eq. (1), invariants, and brute force.  No GPU needed."""
import itertools

import networkx as nx
import numpy as np
import pytest

INT32_MAX = 2 ** 31 - 1


# ----------------------------------------------------------------------------
# An independent statement of the model: positions in the stage order given in
# closed form (not by building the list), the dependency graph made explicit,
# and networkx doing the longest path.
# ----------------------------------------------------------------------------
def _pos_f(w, m):
    return m if m < w else 2 * m - w


def _pos_b(w, M, k):
    return w + 2 * k + 1 if k < M - w else M + k


def build_dag(S, M, t_f, t_b, w, cf, cb):
    """Nodes ('F'|'B', s, m); edge weight = delay + duration of the head node
    (Section 3.1 dependency rules; Section 4.1 / 4.3 stage order)."""
    wc = [min(max(int(x), 0), M - 1) for x in w]
    G = nx.DiGraph()
    dur = {}
    for s in range(S):
        order = [None] * (2 * M)
        for m in range(M):
            order[_pos_f(wc[s], m)] = ("F", s, m)
            order[_pos_b(wc[s], M, m)] = ("B", s, m)
        assert all(o is not None for o in order)
        for m in range(M):
            dur[("F", s, m)] = int(t_f[s])
            dur[("B", s, m)] = int(t_b[s])
        for a, b in zip(order[:-1], order[1:]):
            G.add_edge(a, b, delay=0)
    for s in range(S):
        for m in range(M):
            if s > 0:
                G.add_edge(("F", s - 1, m), ("F", s, m), delay=int(cf[s - 1]))
            if s < S - 1:
                G.add_edge(("B", s + 1, m), ("B", s, m), delay=int(cb[s]))
            else:
                G.add_edge(("F", s, m), ("B", s, m), delay=0)
    for u, v, d in G.edges(data=True):
        d["weight"] = d["delay"] + dur[v]
    for v in list(dur):
        G.add_edge("src", v, delay=0, weight=dur[v])
    return G, dur


def dag_finish_times(G):
    fin = {"src": 0}
    for v in nx.topological_sort(G):
        if v == "src":
            continue
        fin[v] = max(fin[u] + G[u][v]["weight"] for u in G.predecessors(v))
    return fin


def rand_instance(rng, S, M, valid=True, c_hi=200):
    t_f = rng.integers(1, 60, S)
    t_b = rng.integers(1, 90, S)
    cf = rng.integers(0, c_hi, max(S - 1, 0))
    cb = rng.integers(0, c_hi, max(S - 1, 0))
    w = rng.integers(0, M + 1, S)
    if valid:
        w = np.sort(w)[::-1].copy()
    return t_f, t_b, w, cf, cb


# ----------------------------------------------------------------------------
@pytest.mark.parametrize("S,M", [(1, 1), (1, 5), (2, 3), (3, 4), (4, 8), (5, 7), (6, 12)])
def test_every_op_time_equals_dag_longest_path(oracle, S, M):
    rng = np.random.default_rng(100 * S + M)
    for trial in range(12):
        t_f, t_b, w, cf, cb = rand_instance(rng, S, M, valid=True)
        G, dur = build_dag(S, M, t_f, t_b, w, cf, cb)
        assert nx.is_directed_acyclic_graph(G)
        fin = dag_finish_times(G)
        tl = oracle.timeline(S, M, t_f, t_b, w, cf, cb)
        assert tl["completed"]
        assert tl["makespan"] == nx.dag_longest_path_length(G, weight="weight")
        for s in range(S):
            for m in range(M):
                assert tl["fin_f"][s, m] == fin[("F", s, m)], (trial, s, m)
                assert tl["fin_b"][s, m] == fin[("B", s, m)], (trial, s, m)
                assert tl["start_f"][s, m] == fin[("F", s, m)] - t_f[s]
                assert tl["start_b"][s, m] == fin[("B", s, m)] - t_b[s]


@pytest.mark.parametrize("S,M", [(2, 3), (3, 3), (3, 4), (2, 5), (4, 3)])
def test_lemma1_deadlock_iff_not_monotone_full_enumeration(oracle, S, M):
    """Lemma 1: in the fixed-order model a warm-up vector runs to completion iff
    w'_s >= w'_{s+1} for all s (w' = w clamped to [0, M-1]); otherwise the graph
    has a cycle and the simulator must stall.  Also pins the counted in-flight
    peak (w'_s + 1) and the flag byte."""
    rng = np.random.default_rng(7)
    t_f, t_b, _, cf, cb = rand_instance(rng, S, M)
    ws = np.array(list(itertools.product(range(M + 1), repeat=S)), dtype=np.int32).T  # [S, C]
    cap = np.full(S, 2, dtype=np.int32)
    r = oracle.eval_pairs(S, M, t_f, t_b, cap, ws, cf[:, None], cb[:, None], want_peak=True)
    for c in range(ws.shape[1]):
        w = ws[:, c]
        wc = np.minimum(w, M - 1)
        monotone = bool(np.all(wc[:-1] >= wc[1:]))
        G, _ = build_dag(S, M, t_f, t_b, w, cf, cb)
        assert nx.is_directed_acyclic_graph(G) == monotone
        flag = int(r["flag"][0, c])
        assert bool(flag & 2) == (not monotone)
        assert bool(flag & 4) == bool(np.any(wc + 1 > cap))
        assert (flag == 1) == (monotone and not np.any(wc + 1 > cap))
        if monotone:
            assert np.array_equal(r["peak"][:, 0, c], wc + 1)
            assert r["makespan"][0, c] == nx.dag_longest_path_length(G, weight="weight")
        else:
            assert r["makespan"][0, c] == INT32_MAX
            assert np.all(r["bubble"][:, 0, c] == INT32_MAX)


@pytest.mark.parametrize("S,M,tf,tb", [(4, 8, 100, 200), (8, 32, 7, 13), (5, 5, 10, 10), (6, 3, 3, 9), (1, 4, 5, 6)])
def test_closed_form_uniform_1f1b_zero_delay(oracle, S, M, tf, tb):
    """Uniform stage times, plain 1F1B (w_s = S-s-1), no delay:
    makespan = (M+S-1)(t_f+t_b) and every stage idles (S-1)(t_f+t_b)."""
    t_f, t_b = np.full(S, tf), np.full(S, tb)
    w = np.arange(S - 1, -1, -1)
    z = np.zeros(max(S - 1, 0), dtype=np.int32)
    tl = oracle.timeline(S, M, t_f, t_b, w, z, z)
    assert tl["makespan"] == (M + S - 1) * (tf + tb)
    assert np.all(tl["idle"] == (S - 1) * (tf + tb))


def test_single_stage_and_single_microbatch_corners(oracle):
    tl = oracle.timeline(1, 1, [7], [9], [0], [], [])
    assert tl["makespan"] == 16 and tl["idle"][0] == 0 and tl["peak"][0] == 1
    tl = oracle.timeline(1, 6, [7], [9], [3], [], [])
    assert tl["makespan"] == 6 * 16 and tl["idle"][0] == 0 and tl["peak"][0] == 4
    # M = 1, S stages: one forward chain then one backward chain
    S = 4
    t_f, t_b = np.array([3, 5, 7, 11]), np.array([2, 4, 6, 8])
    cf, cb = np.array([10, 20, 30]), np.array([1, 2, 3])
    tl = oracle.timeline(S, 1, t_f, t_b, [5, 3, 1, 0], cf, cb)
    assert tl["makespan"] == t_f.sum() + t_b.sum() + cf.sum() + cb.sum()


def test_gpipe_corner_all_forwards_first(oracle):
    """w_s >= M-1 on every stage (all forwards before any backward), uniform
    times, arbitrary delays: makespan = (M+S-1)(t_f+t_b) + sum of all link delays."""
    rng = np.random.default_rng(3)
    for S, M in [(2, 4), (4, 6), (6, 5)]:
        for _ in range(10):
            tf, tb = int(rng.integers(1, 50)), int(rng.integers(1, 50))
            cf, cb = rng.integers(0, 500, S - 1), rng.integers(0, 500, S - 1)
            tl = oracle.timeline(S, M, np.full(S, tf), np.full(S, tb), np.full(S, M + 3), cf, cb)
            assert tl["makespan"] == (M + S - 1) * (tf + tb) + cf.sum() + cb.sum()


def test_lower_bound_and_identities(oracle):
    """makespan >= critical chain through the last stage; makespan == finish of
    B(0, M-1); accumulated idle gaps == makespan - M (t_f + t_b)."""
    rng = np.random.default_rng(11)
    for _ in range(60):
        S, M = int(rng.integers(2, 7)), int(rng.integers(2, 12))
        t_f, t_b, w, cf, cb = rand_instance(rng, S, M, valid=True, c_hi=400)
        w[S - 1] = 0
        tl = oracle.timeline(S, M, t_f, t_b, w, cf, cb)
        tau = t_f + t_b
        lb = tau[: S - 1].sum() + cf.sum() + cb.sum() + M * tau[S - 1]
        assert tl["makespan"] >= lb
        assert tl["makespan"] == tl["fin_b"][0, M - 1]
        assert np.array_equal(tl["idle"], tl["makespan"] - M * tau)
        # dependencies hold literally (Section 3.1)
        for s in range(S):
            for m in range(M):
                if s > 0:
                    assert tl["start_f"][s, m] >= tl["fin_f"][s - 1, m] + cf[s - 1]
                if s < S - 1:
                    assert tl["start_b"][s, m] >= tl["fin_b"][s + 1, m] + cb[s]
                else:
                    assert tl["start_b"][s, m] >= tl["fin_f"][s, m]


def test_monotone_in_every_delay_and_duration(oracle):
    """Raising any link delay or op duration never lowers a candidate's makespan,
    nor the per-scenario minimum."""
    rng = np.random.default_rng(5)
    for _ in range(25):
        S, M = int(rng.integers(2, 6)), int(rng.integers(2, 10))
        t_f, t_b, _, cf, cb = rand_instance(rng, S, M)
        C = 24
        ws = np.sort(rng.integers(0, M, (S, C)), axis=0)[::-1].astype(np.int32)
        base = oracle.eval_pairs(S, M, t_f, t_b, None, ws, cf[:, None], cb[:, None])["makespan"][0]
        for _ in range(6):
            t_f2, t_b2, cf2, cb2 = t_f.copy(), t_b.copy(), cf.copy(), cb.copy()
            which = rng.integers(0, 4)
            bump = int(rng.integers(1, 300))
            if which == 0:
                cf2[rng.integers(0, S - 1)] += bump
            elif which == 1:
                cb2[rng.integers(0, S - 1)] += bump
            elif which == 2:
                t_f2[rng.integers(0, S)] += bump
            else:
                t_b2[rng.integers(0, S)] += bump
            up = oracle.eval_pairs(S, M, t_f2, t_b2, None, ws, cf2[:, None], cb2[:, None])["makespan"][0]
            assert np.all(up >= base)
            assert up.min() >= base.min()


def _growth(oracle, S, t_f, t_b, w, cf, cb, M0, step, n):
    a = oracle.timeline(S, M0, t_f, t_b, w, cf, cb)["makespan"]
    b = oracle.timeline(S, M0 + n * step, t_f, t_b, w, cf, cb)["makespan"]
    return a, b


@pytest.mark.parametrize("delta", [1, 2, 3, 4])
def test_theorem1_threshold_uniform_times(oracle, delta):
    """Theorem 1 with t_f = t_b = t and one slow link i (delay c both ways):
    c <= (delta-1) t  -> the delay costs a bounded amount, independent of M;
    c >  (delta-1) t  -> every delta+1 further micro-batches cost 4t + 2c
                         (the feasible interval grows from 2 delta t to 2c + 2t),
                         i.e. the extra time grows like M c / (delta + 1)."""
    S, t, link = 4, 10, 1
    t_f = t_b = np.full(S, t)
    w = np.zeros(S, dtype=np.int64)
    for s in range(S - 2, -1, -1):                 # slack `delta` on the slow link, 1 elsewhere
        w[s] = w[s + 1] + (delta if s == link else 1)
    M0 = 40
    for c in range(0, 6 * t + 1, 5):
        cf = np.zeros(S - 1, dtype=np.int64)
        cf[link] = c
        cb = cf.copy()
        z = np.zeros(S - 1, dtype=np.int64)
        a0, b0 = _growth(oracle, S, t_f, t_b, w, z, z, M0, delta + 1, 10)
        a, b = _growth(oracle, S, t_f, t_b, w, cf, cb, M0, delta + 1, 10)
        assert b0 - a0 == 10 * (delta + 1) * 2 * t
        if c <= (delta - 1) * t:
            assert a - a0 == b - b0 == 2 * c            # absorbed: one-off cost only
        else:
            assert b - a == 10 * (4 * t + 2 * c)        # cascading: linear in M
            assert (b - b0) > (a - a0)


def test_eq1_absorption_condition_heterogeneous(oracle):
    """Eq. (1): with non-uniform stage times the delay on link i is absorbed iff
    t_f[i] + t_b[i] + 2 c <= delta_i (t_f[i+1] + t_b[i+1]).  Stage i+1 is made the
    slowest stage so that its period is the pipeline's period when nothing cascades."""
    rng = np.random.default_rng(17)
    S, link = 5, 2
    for _ in range(40):
        t_f = rng.integers(5, 20, S)
        t_b = rng.integers(5, 30, S)
        t_f[link + 1] += 25
        t_b[link + 1] += 35                             # stage link+1 strictly slowest
        tau = t_f + t_b
        delta = int(rng.integers(1, 4))
        w = np.zeros(S, dtype=np.int64)
        for s in range(S - 2, -1, -1):
            w[s] = w[s + 1] + (delta if s == link else 3)   # ample slack on the other links
        c = int(rng.integers(0, 120))
        cf = np.zeros(S - 1, dtype=np.int64)
        cf[link] = c
        cb = cf.copy()
        n, step, M0 = 8, delta + 1, 60
        a, b = _growth(oracle, S, t_f, t_b, w, cf, cb, M0, step, n)
        per_group = (b - a) // n
        assert (b - a) % n == 0
        if tau[link] + 2 * c <= delta * tau[link + 1]:
            assert per_group == step * tau[link + 1]    # no cascading bubbles
        else:
            assert per_group == tau[link] + tau[link + 1] + 2 * c
            assert per_group > step * tau[link + 1]


def test_absorbed_regime_exact_makespan(oracle):
    """Uniform times and Eq. (1) (directional form, c_fwd + c_bwd in place of 2c)
    true on every link: nothing cascades and
    makespan = (M+S-1)(t_f+t_b) + sum of all link delays."""
    rng = np.random.default_rng(23)
    hits = 0
    for _ in range(300):
        S, M = int(rng.integers(2, 7)), int(rng.integers(8, 40))
        tf, tb = int(rng.integers(1, 40)), int(rng.integers(1, 40))
        tau = tf + tb
        d = rng.integers(1, 4, S - 1)
        w = np.concatenate([np.cumsum(d[::-1])[::-1], [0]])
        if w[0] > M - 1:
            continue
        cf = np.array([rng.integers(0, (x - 1) * tau + 1) for x in d])
        cb = np.array([rng.integers(0, (x - 1) * tau - cf[i] + 1) for i, x in enumerate(d)])
        assert np.all(tau + cf + cb <= d * tau)
        tl = oracle.timeline(S, M, np.full(S, tf), np.full(S, tb), w, cf, cb)
        assert tl["makespan"] == (M + S - 1) * tau + cf.sum() + cb.sum()
        hits += 1
    assert hits > 100


@pytest.mark.parametrize("S,M", [(2, 4), (3, 4), (4, 3), (3, 6)])
def test_argmin_brute_force_over_every_warmup_vector(oracle, S, M):
    """best_from_eval against a literal loop over every w in [0, M]^S."""
    rng = np.random.default_rng(31 + S * M)
    t_f, t_b, _, _, _ = rand_instance(rng, S, M)
    K = 5
    cf = rng.integers(0, 300, (S - 1, K))
    cb = rng.integers(0, 300, (S - 1, K))
    cap = rng.integers(2, M + 2, S)
    ws = np.array(list(itertools.product(range(M + 1), repeat=S)), dtype=np.int32).T
    r = oracle.eval_pairs(S, M, t_f, t_b, cap, ws, cf, cb)
    best = oracle.best_from_eval(r["makespan"], r["flag"], r["bubble"])
    for k in range(K):
        bi, bv = -1, INT32_MAX
        for c in range(ws.shape[1]):
            wc = np.minimum(ws[:, c], M - 1)
            if np.any(wc[:-1] < wc[1:]) or np.any(wc + 1 > cap):
                continue
            G, _ = build_dag(S, M, t_f, t_b, ws[:, c], cf[:, k], cb[:, k])
            v = nx.dag_longest_path_length(G, weight="weight")
            if v < bv:
                bi, bv = c, v
        assert best["best_idx"][k] == bi
        assert best["best_makespan"][k] == bv
        if bi >= 0:
            assert np.array_equal(best["best_bubble"][k], bv - M * (t_f + t_b))


def test_no_feasible_candidate_and_histogram(oracle):
    S, M = 3, 4
    t_f, t_b = np.array([5, 6, 7]), np.array([8, 9, 10])
    ws = np.array([[0, 2, 1], [1, 1, 1], [2, 0, 0]], dtype=np.int32)   # cand 0 deadlocks
    cf = cb = np.array([[1, 50], [2, 60]])
    cap_none = np.array([1, 1, 1])                                       # nobody fits
    r = oracle.eval_pairs(S, M, t_f, t_b, cap_none, ws, cf, cb)
    best = oracle.best_from_eval(r["makespan"], r["flag"], r["bubble"])
    assert np.all(best["best_idx"] == -1) and np.all(best["best_makespan"] == INT32_MAX)
    r = oracle.eval_pairs(S, M, t_f, t_b, None, ws, cf, cb)
    assert list(r["flag"][0]) == [2, 1, 1]
    h = oracle.hist_from_eval(r["bubble"], r["flag"], bins=4, shift=5)
    assert h.shape == (S, 4) and np.all(h.sum(axis=1) == 4)
    for s in range(S):
        want = np.zeros(4, dtype=np.uint64)
        for k in range(2):
            for c in (1, 2):
                want[min(3, int(r["bubble"][s, k, c]) >> 5)] += 1
        assert np.array_equal(h[s], want)


def test_pair_list_matches_full_sweep_and_threads_agree(oracle):
    from paper_2504_19232_amd import workloads
    wl = workloads.random_workload(5, S=5, M=9, C=37, K=11)
    full = oracle.eval_workload(wl, threads=1)
    full8 = oracle.eval_workload(wl, threads=8)
    for k in ("makespan", "flag", "bubble"):
        assert np.array_equal(full[k], full8[k])
    pc, ps = workloads.sample_pairs(1, wl.n_cand, wl.n_scen, 200)
    part = oracle.eval_workload(wl, pair_cand=pc, pair_scen=ps)
    assert np.array_equal(part["makespan"], full["makespan"][ps, pc])
    assert np.array_equal(part["flag"], full["flag"][ps, pc])
    assert np.array_equal(part["bubble"], full["bubble"][:, ps, pc])


def test_rejects_negative_times(oracle):
    with pytest.raises(ValueError):
        oracle.timeline(2, 2, [1, -1], [1, 1], [1, 0], [0], [0])
    with pytest.raises(ValueError):
        oracle.timeline(2, 2, [1, 1], [1, 1], [1, 0], [-5], [0])


def test_fb_simulator_agrees_with_the_paper_pinned_fbw_simulator(oracle):
    """Cross-pin: the F/B/W fixed-plan executor (which reproduces the 390 / 400 / 440 ms the paper
    prints, see test_oracle_zb_pins.py) run on a 1F1B-family plan with zero-length W ops must
    give the F/B simulator's makespan and stage idle times."""
    rng = np.random.default_rng(77)
    for _ in range(40):
        S, M = int(rng.integers(1, 7)), int(rng.integers(1, 12))
        t_f, t_b, w, cf, cb = rand_instance(rng, S, M, valid=True, c_hi=300)
        wc = np.minimum(w, M - 1)
        plan = np.zeros((S, 3 * M), dtype=np.int32)
        for s in range(S):
            ops = [None] * (2 * M)
            for m in range(M):
                ops[_pos_f(wc[s], m)] = 0 * M + m
                ops[_pos_b(wc[s], M, m)] = 1 * M + m
            seq = []
            for op in ops:
                seq.append(op)
                if op >= M:
                    seq.append(2 * M + (op - M))          # W(m) right behind B(m), zero length
            plan[s] = seq
        zb = oracle.zb_simulate(S, M, t_f, t_b, np.zeros(S, dtype=np.int32), cf, cb, order=plan)
        tl = oracle.timeline(S, M, t_f, t_b, w, cf, cb)
        assert zb["makespan"] == tl["makespan"]
        assert np.array_equal(zb["idle"], tl["idle"])
        assert np.array_equal(zb["fin"][:, 0, :], tl["fin_f"]) and np.array_equal(zb["fin"][:, 1, :], tl["fin_b"])
