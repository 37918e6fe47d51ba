"""Pins for the ZeroBubble (F / B / W) oracle: the worked example the paper prints, an
explicit dependency graph solved by a library longest-path routine, and invariants."""
import os

import networkx as nx
import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def read_example():
    ex = {"rows": []}
    for line in open(os.path.join(GOLDEN, "paper_zb_example.txt")):
        p = line.split()
        if not p or p[0].startswith("#"):
            continue
        if p[0] in ("S", "N", "t"):
            ex[p[0]] = int(p[1])
        elif p[0] == "x":
            ex["x"] = [int(v) for v in p[1:]]
        elif p[0].startswith("first_backward"):
            ex["b1"] = int(p[1])
        else:
            ex["rows"].append((int(p[0]), int(p[1])))
    return ex


def test_paper_worked_example_390_400_440(oracle):
    """The schedule the selection policy generates without delays must take 390 ms, and that
    same fixed plan executed under 10 / 20 ms on link 0 <-> 1 must take 400 / 440 ms, with the
    first backward of stage 0 starting at 110 ms in the 20 ms case (values printed in the paper)."""
    ex = read_example()
    S, N, t = ex["S"], ex["N"], ex["t"]
    tt = [t] * S
    zero = [0] * (S - 1)
    gen = oracle.zb_simulate(S, N, tt, tt, tt, zero, zero, x=ex["x"])
    assert gen["makespan"] == ex["rows"][0][1] == 390000
    assert gen["start"][S - 1, 0, 0] == (S - 1) * t           # the last stage starts after S-1 forwards upstream
    assert gen["idle"][S - 1] == (S - 1) * t                  # ... and never idles afterwards ("zero bubbles")
    for delay, want in ex["rows"]:
        c = [delay] + [0] * (S - 2)
        r = oracle.zb_simulate(S, N, tt, tt, tt, c, c, order=gen["order"])
        assert r["makespan"] == want, (delay, r["makespan"])
        if delay == 20000:
            assert r["start"][0, 1, 0] == ex["b1"]            # B_1 on stage 0
            assert r["start"][0, 0, 7] == ex["b1"] + t        # F_8 right behind it
    # with its own schedule generated UNDER the delay, the pipeline loses only the delay itself
    for delay in (10000, 20000):
        c = [delay] + [0] * (S - 2)
        assert oracle.zb_simulate(S, N, tt, tt, tt, c, c, x=ex["x"])["makespan"] == 390000 + delay


def zb_dag(S, N, tF, tB, tW, order, cf, cb):
    """Explicit dependency graph of a fixed plan (Section 3.1 rules + the plan's stage order)."""
    dur = lambda ty, i: (tF[i], tB[i], tW[i])[ty]
    G = nx.DiGraph()
    for i in range(S):
        seq = [(int(op) // N, i, int(op) % N) for op in order[i]]
        for a, b in zip(seq[:-1], seq[1:]):
            G.add_edge(a, b, weight=dur(b[0], i))
        for ty, _, m in seq:
            G.add_edge("src", (ty, i, m), weight=dur(ty, i))
            if ty == 0 and i > 0:
                G.add_edge((0, i - 1, m), (0, i, m), weight=cf[i - 1] + dur(0, i))
            if ty == 1:
                if i < S - 1:
                    G.add_edge((1, i + 1, m), (1, i, m), weight=cb[i] + dur(1, i))
                else:
                    G.add_edge((0, i, m), (1, i, m), weight=dur(1, i))
            if ty == 2:
                G.add_edge((1, i, m), (2, i, m), weight=dur(2, i))
    return G


def test_fixed_plan_times_equal_dag_longest_path(oracle):
    rng = np.random.default_rng(4)
    for _ in range(30):
        S, N = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        tF, tB, tW = rng.integers(1, 40, S), rng.integers(1, 40, S), rng.integers(0, 40, S)
        cf, cb = rng.integers(0, 120, max(S - 1, 0)), rng.integers(0, 120, max(S - 1, 0))
        x = np.sort(rng.integers(0, N + 2, S))[::-1]
        gen = oracle.zb_simulate(S, N, tF, tB, tW, cf, cb, x=x)
        assert gen["makespan"] is not None
        # every stage ran each of its 3N ops exactly once
        for i in range(S):
            assert sorted(gen["order"][i]) == list(range(3 * N))
        # replaying the generated plan under the same delays reproduces every time
        rep = oracle.zb_simulate(S, N, tF, tB, tW, cf, cb, order=gen["order"])
        assert rep["makespan"] == gen["makespan"] and np.array_equal(rep["fin"], gen["fin"])
        # ... and under other delays it equals the longest path of the explicit graph
        cf2, cb2 = rng.integers(0, 300, max(S - 1, 0)), rng.integers(0, 300, max(S - 1, 0))
        rep2 = oracle.zb_simulate(S, N, tF, tB, tW, cf2, cb2, order=gen["order"])
        G = zb_dag(S, N, tF, tB, tW, gen["order"], cf2, cb2)
        assert nx.is_directed_acyclic_graph(G)
        assert rep2["makespan"] == nx.dag_longest_path_length(G, weight="weight")
        fin = {"src": 0}
        for v in nx.topological_sort(G):
            if v != "src":
                fin[v] = max(fin[u] + G[u][v]["weight"] for u in G.predecessors(v))
        for (ty, i, m), f in ((k, v) for k, v in fin.items() if k != "src"):
            assert rep2["fin"][i, ty, m] == f


def test_policy_invariants(oracle):
    """Generated schedules obey the policy: the first x_i ops of a stage are forwards (warm-up
    quota), a stage never idles while one of its ops is available, and after the warm-up it
    never runs F or W while a B is available, nor W while an F is available."""
    rng = np.random.default_rng(8)
    for _ in range(25):
        S, N = int(rng.integers(2, 6)), int(rng.integers(2, 10))
        tF, tB, tW = rng.integers(1, 30, S), rng.integers(1, 30, S), rng.integers(1, 30, S)
        cf, cb = rng.integers(0, 90, S - 1), rng.integers(0, 90, S - 1)
        x = np.sort(rng.integers(1, N + 1, S))[::-1]
        g = oracle.zb_simulate(S, N, tF, tB, tW, cf, cb, x=x)
        st, fin, order = g["start"], g["fin"], g["order"]
        for i in range(S):
            assert all(op // N == 0 for op in order[i][: x[i]])
            ready = np.full((3, N), -1, dtype=np.int64)
            ready[0] = 0 if i == 0 else fin[i - 1, 0] + cf[i - 1]
            ready[1] = fin[i, 0] if i == S - 1 else fin[i + 1, 1] + cb[i]
            ready[2] = fin[i, 1]
            assert np.all(st[i] >= ready)
            for pos, op in enumerate(order[i]):
                ty, m = int(op) // N, int(op) % N
                t0 = st[i, ty, m]
                waiting = lambda q: np.any((ready[q] <= t0) & (st[i, q] > t0))
                if pos >= x[i]:
                    if ty != 1:
                        assert not waiting(1)
                    if ty == 2:
                        assert not waiting(0)
                # lowest micro-batch first within a type
                assert not np.any((ready[ty][:m] <= t0) & (st[i, ty][:m] > t0))
            # no idling while something it may run is available
            ends = np.sort(fin[i].ravel())
            starts = np.sort(st[i].ravel())
            for e, s_next in zip(ends[:-1], starts[1:]):
                if s_next > e:
                    for q in range(3):
                        avail = (ready[q] <= e) & (st[i, q] >= s_next)
                        if np.any(avail):
                            # only allowed while the warm-up quota blocks B and W
                            assert q != 0 and np.sum(st[i, 0] < s_next) < x[i]


def test_batch_matches_single(oracle):
    rng = np.random.default_rng(2)
    S, N, C, K = 4, 6, 9, 5
    tF, tB, tW = rng.integers(1, 30, S), rng.integers(1, 30, S), rng.integers(1, 30, S)
    x = np.sort(rng.integers(0, N + 3, (S, C)), axis=0)[::-1].astype(np.int32)
    cf, cb = rng.integers(0, 90, (S - 1, K)), rng.integers(0, 90, (S - 1, K))
    r = oracle.zb_batch(S, N, tF, tB, tW, x, cf, cb)
    for k in range(K):
        for c in range(C):
            one = oracle.zb_simulate(S, N, tF, tB, tW, cf[:, k], cb[:, k], x=x[:, c])
            assert r["makespan"][k, c] == one["makespan"]
            assert np.array_equal(r["idle"][:, k, c], one["idle"])
            assert np.array_equal(one["idle"], one["makespan"] - N * (tF + tB + tW))
